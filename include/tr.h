/*
 * Token Recycling decode step for MI355X (gfx950) — C ABI.
 *
 * One decode step of the method is three calls on one HIP stream:
 *
 *   tr_build_tree         draft: gather the static draft tree from the adjacency matrix
 *   tr_verify_forward     verify: one transformer forward over all tree nodes with tree
 *                         attention, then the per-node top-k over the vocabulary
 *   tr_accept_and_update  accept the longest correct root-to-node path, write every node's
 *                         top-k into the adjacency matrix, compact the accepted K/V
 *
 * Conventions
 *   - Every pointer is tagged [host] or [device] below.  Device pointers must belong to
 *     the HIP device that was current at tr_create.
 *   - Every function returns a tr_status and never throws.  All argument validation is done
 *     on the host before the first HIP call of that function, so each error below can be
 *     provoked without a GPU.
 *   - After tr_create no function allocates device memory; scratch comes from the caller
 *     through the workspace argument (size from tr_workspace_bytes).
 *   - Work is enqueued on the given stream (a hipStream_t passed as void*; NULL = the
 *     default stream).  Nothing synchronises unless stated.
 *   - Calls on one tr_ctx must be issued from one thread at a time.
 *   - Matrices are row-major.  Weight matrices are [out_features, in_features].
 */
#ifndef TR_H
#define TR_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define TR_MAX_NODES 128  /* tree rows including the root                      */
#define TR_PREFILL_ROWS 512 /* prompt rows one ingestion pass takes (packed models) */
#define TR_MAX_LAYERS 32  /* tree layers including the root layer              */
#define TR_MAX_K 32       /* candidates per token (columns of the matrix)      */

typedef struct tr_ctx tr_ctx; /* opaque; owns the adjacency matrix and the device copy of the template */

typedef enum {
  TR_OK = 0,
  TR_EINVAL = -1,    /* NULL pointer, non-positive size, inconsistent shapes, unsupported dtype */
  TR_ETEMPLATE = -2, /* malformed tree template                                                */
  TR_ENOMEM = -3,    /* host or device allocation failed (tr_create only)                      */
  TR_EHIP = -4,      /* a HIP runtime call failed                                              */
  TR_ECAPACITY = -5, /* KV cache or workspace too small for this call                          */
  TR_ESTATE = -6     /* call made in a state that does not allow it                            */
} tr_status;

typedef enum { TR_F32 = 0, TR_BF16 = 1 } tr_dtype;

/*
 * Storage order of the projection and LM-head matrices of a model.
 *   TR_ROW_MAJOR : [out_features, in_features] row-major.
 *   TR_PACKED    : bf16 only; the order the MI355X matrix cores consume directly (written by
 *                  tr_pack_weight): the matrix is cut into tiles of 16 out-features x 32
 *                  in-features, tile (o/16, i/32) stored at ((o/16) * (in/32) + i/32) KiB, and inside
 *                  a tile element (o, i) sits at 16-byte slot (o%16) + 16*((i%32)/8), element i%8.
 *                  Needs out_features % 32 == 0 and in_features % 32 == 0.  The query and key
 *                  projections (wq, wk) are packed by tr_pack_weight_rope instead: their rows are
 *                  first interleaved per head so that the two features a rotary embedding rotates
 *                  together become neighbours.  Queries and cached keys of such a model carry the
 *                  interleaved feature order (the attention dot product is indifferent to it); cached
 *                  values are in natural order.  This is the fast path; row-major models run through
 *                  slower shape-generic kernels.
 * The embedding table and the norm gains are always plain arrays.
 */
typedef enum { TR_ROW_MAJOR = 0, TR_PACKED = 1 } tr_layout;

/*
 * Static draft tree (Section 3.2 "Draft Tree Retrieval", Appendix A.2): the shape is fixed
 * across steps; node i is filled with the rank[i]-th candidate of its parent's token.
 * Nodes are listed layer by layer (breadth-first), root first.  [host], copied at tr_create.
 */
typedef struct {
  int32_t n_nodes;       /* N including the root, 1..TR_MAX_NODES                       */
  int32_t n_layers;      /* D including the root layer, 1..TR_MAX_LAYERS                */
  const int32_t *parent; /* [N]; parent[0] = -1; 0 <= parent[i] < i; depths non-decreasing */
  const int32_t *rank;   /* [N]; rank[0] = -1; 0 <= rank[i] < k; (parent, rank) pairs unique */
} tr_tree_template;

/* Per-layer weights, [device], element type tr_model.dtype. */
typedef struct {
  const void *attn_norm; /* [d_model]                        */
  const void *wq;        /* [n_heads * head_dim, d_model]    */
  const void *wk;        /* [n_kv_heads * head_dim, d_model] */
  const void *wv;        /* [n_kv_heads * head_dim, d_model] */
  const void *wo;        /* [d_model, n_heads * head_dim]    */
  const void *ffn_norm;  /* [d_model]                        */
  const void *w_gate;    /* [d_ffn, d_model]                 */
  const void *w_up;      /* [d_ffn, d_model]                 */
  const void *w_down;    /* [d_model, d_ffn]                 */
} tr_layer;

/*
 * Decoder-only transformer the draft tree is verified with (Section 2.2: one forward pass over
 * the content plus all draft tokens).  The paper uses unmodified Llama-family checkpoints; this
 * is that public architecture: pre-RMSNorm, rotary embedding with half-split pairing
 * (i, i + head_dim/2), grouped-query attention scaled by 1/sqrt(head_dim), SwiGLU FFN, final
 * RMSNorm, untied LM head, no biases.  The struct and the tr_layer array are [host]; the weight
 * pointers inside are [device] and stay owned by the caller.
 */
typedef struct {
  int32_t dtype;  /* tr_dtype of every weight, of the embedding and of the KV cache */
  int32_t layout; /* tr_layout of wq..w_down and lm_head                             */
  int32_t n_layers, d_model, n_heads, n_kv_heads, head_dim, d_ffn, vocab;
  float rms_eps, rope_theta;
  const void *embed;      /* [vocab, d_model] */
  const tr_layer *layers; /* [host] array of n_layers entries */
  const void *final_norm; /* [d_model] */
  const void *lm_head;    /* [vocab, d_model] */
} tr_model;

/*
 * KV cache, owned by the caller, zero-initialised by the caller before first use (stale slots are
 * multiplied by exact zeros, so they must hold finite values).  Positions 0..*d_len-1 are committed
 * (the content so far); tr_verify_forward additionally writes the N tree nodes' keys/values at
 * positions *d_len .. *d_len+N-1, and tr_accept_and_update moves the accepted ones to the front of
 * that range.  Both k and v are [n_layers][n_kv_heads] blocks of capacity * head_dim elements of type
 * dtype; inside a block, element (position p, feature d) sits at
 *   TR_KV_PLAIN : k: p * head_dim + d            v: d * capacity + p   (position-contiguous)
 *   TR_KV_TILED : bf16, head_dim 128, capacity % 32 == 0 only — the operand order of the MI355X
 *                 matrix cores, required by the fast attention kernel:
 *                 k: ((p/16)*4 + d/32)*512 + ((p%16) + 16*((d%32)/8))*8 + d%8
 *                 v: ((p/32)*8 + d/16)*512 + ((d%16) + 16*((p%16)/4))*8 + ((p/16)%2)*4 + p%4
 * len_bound is a host-side upper bound of *d_len kept by the library so that capacity can be
 * checked without reading the device: set both to the same value when (re)initialising.
 */
typedef enum { TR_KV_PLAIN = 0, TR_KV_TILED = 1 } tr_kv_layout;
typedef struct {
  int32_t dtype, layout, n_layers, n_kv_heads, head_dim, capacity;
  void *k;           /* [device] */
  void *v;           /* [device] */
  int32_t *d_len;    /* [device] one int32: committed length L */
  int32_t len_bound; /* [host]   L <= len_bound always          */
} tr_kv;

/* Result of one step, written by tr_accept_and_update. */
typedef struct {
  int32_t n_accepted;             /* a: draft tokens confirmed, 0..D-1                          */
  int32_t n_emitted;              /* a + 1: confirmed drafts plus the model's own next token    */
  int32_t winner;                 /* tree node whose output is that next token                  */
  int32_t next_root;              /* = emitted[a]; root of the next step's tree                 */
  int32_t kv_len;                 /* committed length after the step                            */
  int32_t path[TR_MAX_LAYERS];    /* node indices root..winner (a + 1 valid entries)            */
  int32_t emitted[TR_MAX_LAYERS]; /* the a + 1 new tokens in order                              */
} tr_step_out;

/*
 * Create a context for vocabulary size V and k candidates per token with a static tree.
 * Allocates the adjacency matrix M[V, k] int32 on the current device, initialised to zero
 * (Section 3.1), and the device copy of the template (depths, ancestor bitmasks, layer
 * offsets).  Errors: TR_EINVAL (NULL, V <= 0, k <= 0, k > TR_MAX_K or k > V), TR_ETEMPLATE, TR_ENOMEM,
 * TR_EHIP.  *out is set only on TR_OK and is released with tr_destroy.
 */
tr_status tr_create(int32_t V, int32_t k, const tr_tree_template *tree, tr_ctx **out);
tr_status tr_destroy(tr_ctx *ctx);

/*
 * Variants of the matrix update the paper compares (Section 5.2 "Update Strategies", Appendix A.5, and
 * "Effect of Rejected Tokens", Table 4).  Default: TR_UPDATE_LAST over all nodes.  TR_UPDATE_FIRST lets the
 * first occurrence of a repeated token own the row; | TR_UPDATE_ACCEPTED_ONLY restricts the update to the
 * nodes of the accepted path (first / last then refer to occurrences on that path).  tr_op_matrix_update
 * has no accepted path and ignores TR_UPDATE_ACCEPTED_ONLY.  Errors: TR_EINVAL (NULL, unknown bits).
 */
typedef enum { TR_UPDATE_LAST = 0, TR_UPDATE_FIRST = 1, TR_UPDATE_ACCEPTED_ONLY = 2 } tr_update_mode;
tr_status tr_set_update_mode(tr_ctx *ctx, int32_t mode);

/*
 * Copy the whole matrix from / to [host] memory, int32 [V * k], synchronously (hot start,
 * Section 3.1: the matrix persists across queries and may be saved and restored).
 */
tr_status tr_matrix_load(tr_ctx *ctx, const int32_t *h_M);
tr_status tr_matrix_store(tr_ctx *ctx, int32_t *h_M);

/*
 * Draft-tree retrieval (Section 3.2, Algorithm 1): S[0] = *d_root and, layer by layer,
 * S[i] = M[S[parent[i]], rank[i]].  d_root [device] one int32 in [0, V); d_S [device] int32 [N],
 * the merged sequence in breadth-first order.  A root, or a stored candidate, outside [0, V) is
 * clamped into range by the kernel (no error is reported from device code).
 */
tr_status tr_build_tree(tr_ctx *ctx, const int32_t *d_root, int32_t *d_S, void *stream);

/*
 * Repack one row-major bf16 matrix d_src [out_f, in_f] into TR_PACKED order at d_dst (same size,
 * must not overlap), on the stream.  Errors: TR_EINVAL (NULL, sizes not multiples of 32).
 */
tr_status tr_pack_weight(const void *d_src, void *d_dst, int32_t out_f, int32_t in_f, void *stream);

/*
 * The same for a query or key projection (Section 2.2: the verification forward is a Llama-style
 * decoder whose attention uses rotary position embedding with half-split pairing): packed row
 * h*head_dim + 2j + b takes source row h*head_dim + j + b*head_dim/2 (b = 0, 1), so that the projection
 * kernel can rotate a pair inside one lane and write queries and keys straight from its epilogue.
 * Errors as tr_pack_weight, plus TR_EINVAL if head_dim is not a positive multiple of 4 dividing out_f.
 */
tr_status tr_pack_weight_rope(const void *d_src, void *d_dst, int32_t out_f, int32_t in_f,
                              int32_t head_dim, void *stream);

/*
 * Launch plan of one packed projection (diagnostic; touches no GPU).  For n_rows activation rows
 * (tree nodes, Section 2.2: all nodes of the draft tree go through the model in one forward) and a
 * weight of [out_f, in_f], reports what tr_verify_forward would launch: plan[0] = most 16-row weight
 * tiles one workgroup owns (gate/up tile pairs when fused_pair != 0, where out_f counts one of the two
 * matrices), plan[1] = workgroups per split of the input dimension, plan[2] = splits of the input
 * dimension (1 .. max_splits; always 1 when fused_pair).  plan is [host], 3 values.
 * TR_EINVAL for null plan, max_splits < 1, or a shape the packed kernels do not take (n_rows outside
 * 1..TR_MAX_NODES, in_f or out_f not a multiple of 32).
 */
tr_status tr_plan_projection(int32_t n_rows, int32_t in_f, int32_t out_f, int32_t fused_pair,
                             int32_t max_splits, int32_t *plan);

/*
 * Launch plan of the tree-attention kernel (Section 2.2 "Tree Attention") for n_heads query heads over
 * n_kv_heads K/V heads, n_nodes tree nodes and a host bound len_bound on committed length + tree nodes
 * (diagnostic; touches no GPU): plan[0] = query heads one workgroup serves (heads sharing a K/V head
 * share its staged tiles), plan[1] = key-axis splits, or 0 for the one-launch form short sequences take (one
 * workgroup per query head and tile of 16 nodes, its waves splitting the keys, no merge pass).  plan is
 * [host], 2 values.  TR_EINVAL for null
 * plan, n_kv_heads < 1, n_heads not a positive multiple of n_kv_heads, n_nodes outside 1..TR_MAX_NODES
 * or len_bound < 1.
 */
tr_status tr_plan_attention(int32_t n_heads, int32_t n_kv_heads, int32_t n_nodes, int32_t len_bound,
                            int32_t *plan);

/* Bytes of [device] workspace tr_verify_forward / tr_prefill need for this model (256-aligned). */
tr_status tr_workspace_bytes(const tr_ctx *ctx, const tr_model *model, size_t *bytes);

/*
 * Verification forward (Section 2.2 "Guess and Verify" and "Tree Attention"): runs the N tokens
 * d_S through the model in one pass.  Node i sits at position L + depth(i) and attends to the
 * committed positions 0..L-1 and to its own ancestors and itself — nothing else, exactly.
 * Writes the nodes' keys/values to cache positions L..L+N-1, the logits to d_logits if it is not
 * NULL ([device] float32 [N, vocab]), and the per-node candidates argtopk (Section 2.1) to
 * d_topk ([device] int32 [N, k]): indices of the k largest logits, largest first, equal values
 * ordered by increasing index (Appendix A.1 tie rule), -0 equal to +0.
 * Errors: TR_EINVAL (NULL, model/cache/ctx shapes disagree, unsupported shape), TR_ECAPACITY
 * (kv->len_bound + N > capacity, or workspace too small), TR_EHIP.
 */
tr_status tr_verify_forward(tr_ctx *ctx, const tr_model *model, tr_kv *kv, const int32_t *d_S,
                            float *d_logits, int32_t *d_topk, void *d_workspace,
                            size_t workspace_bytes, void *stream);

/*
 * Accept and update (Section 3.3 "Verification and Update").  With out[i] = d_topk[i, 0]:
 * node i is correct when every draft token on its root-to-node path equals the output at that
 * token's parent; the deepest correct node wins (smallest index among equals).  Then
 *   - emitted = the winner's path tokens after the root, then out[winner];
 *   - M[S[i], :] = d_topk[i, :] for ALL N nodes (accepted, rejected and the root); a token that
 *     occurs several times keeps the candidates of its last occurrence (Appendix A.5 "Last",
 *     one of the outcomes the paper's unordered update can produce);
 *   - the path nodes' keys/values move to cache positions L..L+a and *kv->d_len becomes L+a+1.
 * d_out [device] receives the result.  If h_out is not NULL ([host]) the result is also copied
 * there and the stream is synchronised; kv->len_bound then becomes exact, otherwise it grows
 * by the tree depth.  Errors: TR_EINVAL, TR_ECAPACITY, TR_EHIP.
 */
tr_status tr_accept_and_update(tr_ctx *ctx, tr_kv *kv, const int32_t *d_S, const int32_t *d_topk,
                               tr_step_out *d_out, tr_step_out *h_out, void *stream);

/*
 * Temperature sampling (Section 5.3 "Temperature Sampling").  The paper reports results under sampling
 * without stating the rule; the reading taken here: the token the model emits at a node is drawn from
 * softmax(logits / T) instead of taken as the argmax, a draft is correct when it equals the token drawn
 * at its parent (the chain rule of Section 2.2 unchanged), and the matrix still stores the top-k of the
 * logits.  The draw is the Gumbel-max form with noise the caller supplies per sequence position:
 *
 *   tr_op_sample: d_tokens[i] = argmax_j ( d_logits[i][j] * inv_temperature
 *                                          + d_noise[(L + depth(i)) - noise_pos0][j] ),
 *     ties to the smallest j, for the N nodes of the context's tree; the multiply and the add are
 *     two separately rounded float32 operations.  d_logits [device] float32 [N, V] as written by
 *     tr_verify_forward; d_noise [device] float32 [noise_rows, V], row r holding the noise of
 *     sequence position noise_pos0 + r (standard Gumbel values give a draw from softmax(logits/T);
 *     zeros give the greedy rule); d_tokens [device] int32 [N].  Call it between tr_verify_forward
 *     and the accept call of the same step (L must not have moved).  Keying the noise by position
 *     makes a tree node and a plain one-token step at the same position draw the same token, so a
 *     run under sampling emits exactly the sequence plain sampling would.
 *     Errors: TR_EINVAL (NULL, noise_pos0 < 0, noise_rows <= 0, inv_temperature not positive and
 *     finite), TR_ECAPACITY (the table does not reach kv->len_bound + n_layers), TR_EHIP.  A position
 *     below noise_pos0 cannot be detected on the host (L lives on the device): the kernel then
 *     reads the table's first row.
 *   tr_accept_and_update_sampled: tr_accept_and_update with d_tokens [device] int32 [N] in the place
 *     of the first top-k column as "the token the model emits at node i".  Errors as there, plus
 *     TR_EINVAL for a NULL d_tokens.
 */
tr_status tr_op_sample(tr_ctx *ctx, const tr_kv *kv, const float *d_logits, const float *d_noise,
                       int32_t noise_pos0, int32_t noise_rows, float inv_temperature,
                       int32_t *d_tokens, void *stream);
tr_status tr_accept_and_update_sampled(tr_ctx *ctx, tr_kv *kv, const int32_t *d_S,
                                       const int32_t *d_topk, const int32_t *d_tokens,
                                       tr_step_out *d_out, tr_step_out *h_out_or_null, void *stream);

/*
 * Prompt ingestion: runs d_tokens [device] int32 [n_tokens] causally after the committed prefix
 * (a chain is a tree whose node i has ancestors 0..i), commits their keys/values and advances
 * *kv->d_len and kv->len_bound by n_tokens.  No logits, no matrix update (the paper updates M only
 * from decoding steps, Section 3.3).  Packed bf16 models with a tiled cache take TR_PREFILL_ROWS
 * tokens per pass (a projection kernel of its own reads each layer's weights once per pass; the
 * tree-attention kernels run per block of TR_MAX_NODES rows; the last layer stops after its K/V
 * are cached); all other models, and what is left after the full passes when it is at most
 * TR_MAX_NODES tokens, go through the decode-step kernels TR_MAX_NODES tokens at a time.  Same
 * arithmetic per token either way.  Errors: TR_EINVAL (NULL, n_tokens < 0, model / cache
 * mismatch), TR_ECAPACITY (kv->len_bound + n_tokens beyond the capacity, workspace smaller than
 * tr_workspace_bytes), TR_EHIP.  n_tokens == 0 is a no-op.
 */
tr_status tr_prefill(tr_ctx *ctx, const tr_model *model, tr_kv *kv, const int32_t *d_tokens,
                     int32_t n_tokens, void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * Single operations of the step, exposed for kernel-level parity tests and microbenchmarks.
 *
 * tr_op_topk: argtopk of each of n_rows rows of d_logits ([device], dtype f32 or bf16,
 *   [n_rows, V] with V the context's vocabulary) into d_topk [device] int32 [n_rows, k].
 * tr_op_matrix_update: the M scatter of tr_accept_and_update alone, all N nodes, last wins.
 * tr_op_tree_attention: the attention of one layer.  d_q [device] [N, n_heads, head_dim]
 *   (already rotated), cache layer `layer` of kv holding L committed positions plus the N tree
 *   nodes' keys/values at L..L+N-1; d_out [device] [N, n_heads, head_dim]; element type kv->dtype.
 * tr_op_linear: y[n_rows, out_f] (float32) = x[n_rows, in_f] * w[out_f, in_f]^T, x row-major and w
 *   row-major or packed (layout), both of element type dtype.  With TR_PACKED the call goes through
 *   the kernel the projections use (x is rearranged into the workspace first; `splits` partial sums
 *   over in_f are added up in order); with TR_ROW_MAJOR through the generic kernel (splits ignored).
 *   n_rows is 1..TR_MAX_NODES; with TR_PACKED up to TR_PREFILL_ROWS, where more than TR_MAX_NODES rows go
 *   through the kernel that prompt ingestion uses (in_f >= 64; it splits over in_f at most `splits` times,
 *   fewer when the launch fills the chip without).
 */
tr_status tr_op_topk(tr_ctx *ctx, const void *d_logits, int32_t dtype, int32_t n_rows,
                     int32_t *d_topk, void *stream);
tr_status tr_op_matrix_update(tr_ctx *ctx, const int32_t *d_S, const int32_t *d_topk, void *stream);
tr_status tr_op_tree_attention(tr_ctx *ctx, const tr_kv *kv, int32_t layer, int32_t n_heads,
                               const void *d_q, void *d_out, void *d_workspace,
                               size_t workspace_bytes, void *stream);
tr_status tr_op_linear(tr_ctx *ctx, const void *d_x, const void *d_w, int32_t dtype, int32_t layout,
                       int32_t n_rows, int32_t in_f, int32_t out_f, int32_t splits, float *d_y,
                       void *d_workspace, size_t workspace_bytes, void *stream);

/*
 * tr_op_topk for callers that cannot allocate device memory and therefore hold no context (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same kernels, with
 * their candidate scratch in a device array that is part of the library image (1 MiB per GPU, held
 * until the process ends) instead of context-owned memory.  Allocates nothing, on the host or the
 * device.  Limits: n_rows <= TR_MAX_NODES, 8 <= V <= 131072, k <= 8; beyond them TR_ECAPACITY
 * (TR_EINVAL for NULL pointers, an unknown dtype, n_rows < 0, V <= 0, k <= 0 or k > V).  Arguments as
 * tr_op_topk, with V and k given explicitly.  All calls on one GPU share that GPU's array: calls
 * that overlap in time on one GPU (different streams or threads) race and must be serialised by
 * the caller; consecutive calls on one stream are safe.
 */
tr_status tr_op_topk_static(const void *d_logits, int32_t dtype, int32_t n_rows, int32_t V, int32_t k,
                            int32_t *d_topk, void *stream);

/*
 * Measurement aid: one plain streaming pass over `bytes` (multiple of 16) of [device] memory with the
 * same load instructions the weight-streaming kernels use — read-only if d_dst is NULL, else a copy
 * to d_dst.  Gives the achievable HBM streaming rate on the machine at hand and a kernel of known
 * traffic to calibrate hardware byte counters against.
 */
tr_status tr_op_stream(const void *d_src, void *d_dst, size_t bytes, void *stream);

/*
 * Per-kernel timing for the time-allocation breakdown (the paper's Figure 6 reports the same
 * split: retrieval / model forward / verification / update).  While enabled, every kernel the
 * step calls launch carries a start and a stop event tied to that dispatch, so an entry's time is
 * the kernels' own execution time (launch latency and the gaps between kernels are not in it);
 * tr_profile_read synchronises the device, sums the times per kernel class, returns up to
 * max_entries entries ([host]) and resets the counters.  Enabling allocates the event pool (the
 * only allocation after tr_create); kernels beyond the pool are launched untimed.
 */
typedef struct {
  char name[24];
  int32_t launches;
  double ms;            /* total elapsed over those launches */
} tr_profile_entry;
tr_status tr_profile_enable(tr_ctx *ctx, int32_t enable);
tr_status tr_profile_read(tr_ctx *ctx, tr_profile_entry *h_entries, int32_t max_entries,
                          int32_t *n_entries);

/* Static, never NULL. */
const char *tr_strerror(tr_status status);

#ifdef __cplusplus
}
#endif
#endif /* TR_H */
