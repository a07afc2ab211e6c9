// Integer kernels of the Token Recycling step: draft-tree gather, per-row top-k, greedy accept,
// adjacency-matrix scatter and KV compaction.  All single-workgroup or tiny: the work is a few
// KB of dependent L2 accesses, so each kernel is shaped to be one launch with no host round trip.
#include "tr_internal.h"

namespace tr {

// ---------------------------------------------------------------------------------------------
// Draft-tree retrieval (Section 3.2, Algorithm 1).  One workgroup; the tree lives in LDS and the
// D-1 dependent gather rounds are separated by workgroup barriers.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(TR_MAX_NODES) void k_build_tree(const int32_t *__restrict__ M, int32_t V,
                                                             int32_t k, TreeDev t,
                                                             const int32_t *__restrict__ d_root,
                                                             int32_t *__restrict__ S) {
  __shared__ int32_t s[TR_MAX_NODES];
  const int i = threadIdx.x;
  const bool live = i < t.n_nodes;
  const int par = live ? t.parent[i] : -1;
  const int rk = live ? t.rank[i] : 0;
  const int dep = live ? t.depth[i] : -1;
  if (i == 0) {
    int r = *d_root;
    s[0] = r < 0 ? 0 : (r >= V ? V - 1 : r);
  }
  for (int d = 1; d < t.n_layers; ++d) {
    __syncthreads();
    if (dep == d) s[i] = M[(size_t)s[par] * k + rk];
  }
  __syncthreads();
  if (live) S[i] = s[i];
}

hipError_t launch_build_tree(const tr_ctx *c, const int32_t *d_root, int32_t *d_S, hipStream_t st) {
  hipLaunchKernelGGL(k_build_tree, dim3(1), dim3(TR_MAX_NODES), 0, st, c->d_M, c->V, c->k, c->tree,
                     d_root, d_S);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// argtopk (Section 2.1): one workgroup per row, k selection passes.  Pass p finds the first
// element, in the total order (value descending, index ascending), that comes strictly after the
// winner of pass p-1.  Exact for ties and for -0 == +0; no per-thread candidate lists.
// ---------------------------------------------------------------------------------------------
struct Cand {
  float v;
  int32_t i;
};
__device__ inline bool before(const Cand &a, const Cand &b) { // a strictly precedes b
  return a.v > b.v || (a.v == b.v && a.i < b.i);
}

constexpr int TOPK_THREADS = 512;

template <typename T>
__global__ __launch_bounds__(TOPK_THREADS) void k_topk(const T *__restrict__ logits, int32_t V, int32_t k,
                                                        int32_t *__restrict__ out) {
  __shared__ Cand red[TOPK_THREADS / 64];
  __shared__ Cand winner;
  const T *row = logits + (size_t)blockIdx.x * V;
  const int tid = threadIdx.x;
  Cand prev;
  prev.v = __builtin_inff();
  prev.i = -1; // precedes every real element
  for (int p = 0; p < k; ++p) {
    Cand best;
    best.v = -__builtin_inff();
    best.i = 0x7FFFFFFF; // follows every real element
    for (int j = tid; j < V; j += TOPK_THREADS) {
      Cand e;
      e.v = to_f32<T>(row[j]);
      e.i = j;
      if (before(prev, e) && before(e, best)) best = e;
    }
    for (int off = 32; off > 0; off >>= 1) {
      Cand o;
      o.v = __shfl_xor(best.v, off);
      o.i = __shfl_xor(best.i, off);
      if (before(o, best)) best = o;
    }
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    if (tid == 0) {
      Cand b = red[0];
      for (int w = 1; w < TOPK_THREADS / 64; ++w)
        if (before(red[w], b)) b = red[w];
      winner = b;
      out[(size_t)blockIdx.x * k + p] = b.i;
    }
    __syncthreads();
    prev = winner;
  }
}

// Two-stage variant for k <= 8.  Stage 1, grid (row, segment): the row is cut into TOPK_SEGS segments;
// every thread loads its (at most TOPK_PER_THREAD) elements of the segment at once, keeps them sorted in
// registers, and k rounds of a workgroup-wide "best head of list" write the segment's k best candidates.
// Stage 2, one wave per row: the TOPK_SEGS * k candidates are merged the same way.  Both stages use the
// total order of k_topk, so ties resolve identically.
constexpr int TOPK_SEGS = 8;
constexpr int TOPK1_THREADS = 256;
constexpr int TOPK_PER_THREAD = 8; // registers per thread; longer segments loop

__device__ inline void insert8(Cand (&l)[8], const Cand &e) {
  if (before(e, l[7])) {
    bool placed = false;
#pragma unroll
    for (int p = 7; p >= 0; --p) {
      if (!placed) {
        if (p > 0 && before(e, l[p - 1])) {
          l[p] = l[p - 1];
        } else {
          l[p] = e;
          placed = true;
        }
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(TOPK1_THREADS) void k_topk_stage1(const T *__restrict__ logits, int32_t V, int32_t k,
                                                                Cand *__restrict__ cand) {
  __shared__ Cand red[TOPK1_THREADS / 64];
  const int rowi = blockIdx.x, seg = blockIdx.y, tid = threadIdx.x;
  const T *row = logits + (size_t)rowi * V;
  const int seg_len = (V + TOPK_SEGS - 1) / TOPK_SEGS;
  const int lo = seg * seg_len;
  const int hi = lo + seg_len < V ? lo + seg_len : V;
  Cand l[8];
#pragma unroll
  for (int p = 0; p < 8; ++p) {
    l[p].v = -__builtin_inff();
    l[p].i = 0x7FFFFFFF; // sentinel: after every real element
  }
  for (int j0 = lo + tid; j0 < hi; j0 += TOPK_PER_THREAD * TOPK1_THREADS) {
    float batch[TOPK_PER_THREAD];
#pragma unroll
    for (int b = 0; b < TOPK_PER_THREAD; ++b) {
      const int j = j0 + b * TOPK1_THREADS;
      batch[b] = j < hi ? to_f32<T>(row[j]) : -__builtin_inff();
    }
#pragma unroll
    for (int b = 0; b < TOPK_PER_THREAD; ++b) {
      Cand e;
      e.v = batch[b];
      e.i = j0 + b * TOPK1_THREADS;
      if (e.i < hi) insert8(l, e);
    }
  }
  for (int p = 0; p < k; ++p) {
    Cand best = l[0];
    for (int off = 32; off > 0; off >>= 1) {
      Cand o;
      o.v = __shfl_xor(best.v, off);
      o.i = __shfl_xor(best.i, off);
      if (before(o, best)) best = o;
    }
    if ((tid & 63) == 0) red[tid >> 6] = best;
    __syncthreads();
    Cand b = red[0];
#pragma unroll
    for (int w = 1; w < TOPK1_THREADS / 64; ++w)
      if (before(red[w], b)) b = red[w];
    if (tid == 0) cand[((size_t)rowi * TOPK_SEGS + seg) * 8 + p] = b;
    // the owner of the winning element pops it (real indices are unique; sentinels never need popping)
    if (l[0].i == b.i && b.i != 0x7FFFFFFF) {
#pragma unroll
      for (int q = 0; q < 7; ++q) l[q] = l[q + 1];
      l[7].v = -__builtin_inff();
      l[7].i = 0x7FFFFFFF;
    }
    __syncthreads();
  }
}

__global__ __launch_bounds__(64) void k_topk_stage2(const Cand *__restrict__ cand, int32_t k, int32_t *__restrict__ out) {
  const int rowi = blockIdx.x, lane = threadIdx.x;
  // lane = segment * 8 + rank; ranks >= k were not written by stage 1
  Cand mine = cand[(size_t)rowi * TOPK_SEGS * 8 + lane];
  if ((lane & 7) >= k) {
    mine.v = -__builtin_inff();
    mine.i = 0x7FFFFFFF;
  }
  for (int p = 0; p < k; ++p) {
    Cand best = mine;
    for (int off = 32; off > 0; off >>= 1) {
      Cand o;
      o.v = __shfl_xor(best.v, off);
      o.i = __shfl_xor(best.i, off);
      if (before(o, best)) best = o;
    }
    if (lane == 0) out[(size_t)rowi * k + p] = best.i;
    if (mine.i == best.i) {
      mine.v = -__builtin_inff();
      mine.i = 0x7FFFFFFF;
    }
  }
}

hipError_t launch_topk(const void *logits, int32_t dtype, int32_t rows, int32_t V, int32_t k, int32_t *d_topk,
                       void *d_cand, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  const size_t esz = dtype_size(dtype);
  if (k <= 8 && V >= TOPK_SEGS * k && d_cand != nullptr) {
    for (int r0 = 0; r0 < rows; r0 += TR_MAX_NODES) { // the candidate scratch holds TR_MAX_NODES rows
      const int nr = rows - r0 < TR_MAX_NODES ? rows - r0 : TR_MAX_NODES;
      const char *src = (const char *)logits + (size_t)r0 * V * esz;
      if (dtype == TR_BF16)
        hipLaunchKernelGGL(k_topk_stage1<bf16_t>, dim3(nr, TOPK_SEGS), dim3(TOPK1_THREADS), 0, st, (const bf16_t *)src, V,
                           k, (Cand *)d_cand);
      else
        hipLaunchKernelGGL(k_topk_stage1<float>, dim3(nr, TOPK_SEGS), dim3(TOPK1_THREADS), 0, st, (const float *)src, V,
                           k, (Cand *)d_cand);
      hipLaunchKernelGGL(k_topk_stage2, dim3(nr), dim3(64), 0, st, (const Cand *)d_cand, k, d_topk + (size_t)r0 * k);
    }
    return hipGetLastError();
  }
  if (dtype == TR_BF16)
    hipLaunchKernelGGL(k_topk<bf16_t>, dim3(rows), dim3(TOPK_THREADS), 0, st, (const bf16_t *)logits, V, k, d_topk);
  else
    hipLaunchKernelGGL(k_topk<float>, dim3(rows), dim3(TOPK_THREADS), 0, st, (const float *)logits, V, k, d_topk);
  return hipGetLastError();
}

size_t topk_scratch_bytes() { return (size_t)TR_MAX_NODES * TOPK_SEGS * 8 * sizeof(Cand); }

// ---------------------------------------------------------------------------------------------
// Matrix update (Section 3.3): M[S[i], :] = topk[i, :] for every node.  A token that occurs more
// than once is written by its last occurrence only (Appendix A.5 "Last"), which makes the result
// independent of thread scheduling.
// ---------------------------------------------------------------------------------------------
// mode: TR_UPDATE_LAST / TR_UPDATE_FIRST (which occurrence of a repeated token owns the row), optionally
// | TR_UPDATE_ACCEPTED_ONLY (only nodes on the accepted path are eligible, e0/e1 = their bit mask).
__device__ inline void scatter_rows(int32_t *__restrict__ M, int32_t k, int n_nodes, const int32_t *sS,
                                    const int32_t *__restrict__ topk, int i, int mode, uint64_t e0, uint64_t e1) {
  if (i >= n_nodes) return;
  const bool restricted = (mode & TR_UPDATE_ACCEPTED_ONLY) != 0;
  auto eligible = [&](int j) { return !restricted || ((j < 64 ? (e0 >> j) : (e1 >> (j - 64))) & 1ull); };
  if (!eligible(i)) return;
  const int tok = sS[i];
  if ((mode & 1) == TR_UPDATE_FIRST) {
    for (int j = 0; j < i; ++j)
      if (sS[j] == tok && eligible(j)) return; // an earlier occurrence owns the row
  } else {
    for (int j = i + 1; j < n_nodes; ++j)
      if (sS[j] == tok && eligible(j)) return; // a later occurrence owns the row
  }
  for (int c = 0; c < k; ++c) M[(size_t)tok * k + c] = topk[(size_t)i * k + c];
}

__global__ __launch_bounds__(TR_MAX_NODES) void k_matrix_update(int32_t *__restrict__ M, int32_t V, int32_t k,
                                                                int32_t n_nodes, const int32_t *__restrict__ S,
                                                                const int32_t *__restrict__ topk, int32_t mode) {
  __shared__ int32_t sS[TR_MAX_NODES];
  const int i = threadIdx.x;
  if (i < n_nodes) {
    int t = S[i];
    sS[i] = t < 0 ? 0 : (t >= V ? V - 1 : t);
  }
  __syncthreads();
  scatter_rows(M, k, n_nodes, sS, topk, i, mode & 1, 0ull, 0ull); // no path here: every node is eligible
}

hipError_t launch_matrix_update(const tr_ctx *c, const int32_t *d_S, const int32_t *d_topk, hipStream_t st) {
  hipLaunchKernelGGL(k_matrix_update, dim3(1), dim3(TR_MAX_NODES), 0, st, c->d_M, c->V, c->k,
                     c->tree.n_nodes, d_S, d_topk, c->update_mode);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Greedy accept + matrix update in one workgroup (Section 3.3 with the chain rule of Section 2.2).
// match bit i  = draft token i equals the model output at its parent (root: always)
// node i is ok = every bit of its ancestor mask is a match bit
// winner       = deepest ok node, smallest index among equals
// The kernel also publishes the committed length before the step (step_L) and advances *d_len, so
// the compaction kernel that follows works from step_L and needs no further bookkeeping launch.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(TR_MAX_NODES) void k_accept_update(int32_t *__restrict__ M, int32_t V, int32_t k,
                                                                TreeDev t, const int32_t *__restrict__ S,
                                                                const int32_t *__restrict__ topk,
                                                                const int32_t *__restrict__ tokens,
                                                                int32_t *__restrict__ d_len,
                                                                int32_t *__restrict__ step_L,
                                                                tr_step_out *__restrict__ out, int32_t mode) {
  __shared__ int32_t sS[TR_MAX_NODES];
  __shared__ int32_t sOut[TR_MAX_NODES];
  __shared__ uint64_t mbits[2];
  __shared__ int32_t best_key;
  const int i = threadIdx.x;
  const bool live = i < t.n_nodes;
  if (i == 0) best_key = -1;
  if (live) {
    int tk = S[i];
    sS[i] = tk < 0 ? 0 : (tk >= V ? V - 1 : tk);
    // the token the model emits at node i: its argmax, or the caller's draw under temperature sampling
    int ot = tokens != nullptr ? tokens[i] : topk[(size_t)i * k];
    sOut[i] = ot < 0 ? 0 : (ot >= V ? V - 1 : ot);
  }
  __syncthreads();
  const bool match = live && (i == 0 || sS[i] == sOut[t.parent[i]]);
  const uint64_t ballot = __ballot(match);
  if ((i & 63) == 0) mbits[i >> 6] = ballot;
  __syncthreads();
  if (live) {
    const uint64_t a0 = t.anc[2 * i], a1 = t.anc[2 * i + 1];
    const bool ok = ((mbits[0] & a0) == a0) && ((mbits[1] & a1) == a1);
    if (ok) atomicMax(&best_key, t.depth[i] * 256 + (255 - i));
  }
  __syncthreads();
  if (i == 0) {
    const int w = 255 - (best_key & 255);
    const int a = best_key >> 8;
    uint64_t a0 = t.anc[2 * w], a1 = t.anc[2 * w + 1];
    int cnt = 0;
    // ancestors in increasing index order are the path root..winner (breadth-first numbering)
    for (int j = 0; j < t.n_nodes; ++j) {
      const bool on = j < 64 ? ((a0 >> j) & 1) : ((a1 >> (j - 64)) & 1);
      if (on) {
        out->path[cnt] = j;
        if (cnt > 0) out->emitted[cnt - 1] = sS[j];
        ++cnt;
      }
    }
    const int bonus = sOut[w];
    out->emitted[a] = bonus;
    for (int j = cnt; j < TR_MAX_LAYERS; ++j) {
      out->path[j] = -1;
      out->emitted[j] = -1;
    }
    out->n_accepted = a;
    out->n_emitted = a + 1;
    out->winner = w;
    out->next_root = bonus;
    const int L = *d_len;
    *step_L = L;
    *d_len = L + a + 1;
    out->kv_len = L + a + 1;
  }
  // best_key is final since the barrier above; every thread derives the winner's path mask from it
  const int win = 255 - (best_key & 255);
  scatter_rows(M, k, t.n_nodes, sS, topk, i, mode, t.anc[2 * win], t.anc[2 * win + 1]);
}

// ---------------------------------------------------------------------------------------------
// KV compaction: the accepted path's keys/values (written by the forward at L + node index) move
// to L + 0..a.  One workgroup per (layer, kv head); all sources are staged in LDS before any
// destination is written, so overlapping source/destination positions are safe.
//   K: [layers][Hkv][cap][hd]   V: [layers][Hkv][hd][cap]
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_compact_kv(T *__restrict__ K, T *__restrict__ Vt, int32_t cap, int32_t hd,
                                                    int32_t tiled, const int32_t *__restrict__ step_L,
                                                    const tr_step_out *__restrict__ out) {
  extern __shared__ unsigned char smem_raw[];
  T *sk = reinterpret_cast<T *>(smem_raw);          // [a+1][hd]
  const int a = out->n_accepted;
  if (a == 0) return;                                 // root already sits at L
  T *sv = sk + (size_t)TR_MAX_LAYERS * hd;           // [a+1][hd]
  const int L = *step_L;
  const size_t blk = blockIdx.x;                     // layer * Hkv + head
  T *Kb = K + blk * (size_t)cap * hd;
  T *Vb = Vt + blk * (size_t)hd * cap;
  const int total = (a + 1) * hd;
  for (int e = threadIdx.x; e < total; e += blockDim.x) {
    const int i = e / hd, d = e - i * hd;
    const int src = L + out->path[i];
    sk[e] = Kb[tiled ? kv_k_index(src, d) : (size_t)src * hd + d];
    sv[e] = Vb[tiled ? kv_v_index(src, d) : (size_t)d * cap + src];
  }
  __syncthreads();
  for (int e = threadIdx.x; e < total; e += blockDim.x) {
    const int i = e / hd, d = e - i * hd;
    const int dst = L + i;
    Kb[tiled ? kv_k_index(dst, d) : (size_t)dst * hd + d] = sk[e];
    Vb[tiled ? kv_v_index(dst, d) : (size_t)d * cap + dst] = sv[e];
  }
}

// ---------------------------------------------------------------------------------------------
// Temperature sampling (Section 5.3): the token drawn at node i is
//   argmax_j ( logits[i][j] * inv_t + noise[L + depth(i) - pos0][j] ),   ties to the smallest j,
// i.e. a draw from softmax(logits / T) when the noise is standard Gumbel.  The two float32 operations
// are kept separate (no fused multiply-add): they decide an integer, and whoever repeats them rounds
// the same way.  One workgroup per node.
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(256) void k_sample_tokens(const float *__restrict__ logits, const float *__restrict__ noise,
                                                       int32_t V, int32_t pos0, int32_t noise_rows, float inv_t,
                                                       const int32_t *__restrict__ depth,
                                                       const int32_t *__restrict__ d_len, int32_t *__restrict__ tokens) {
  __shared__ float sv[256];
  __shared__ int32_t si[256];
  const int i = blockIdx.x;
  int row = *d_len + depth[i] - pos0;
  row = row < 0 ? 0 : (row >= noise_rows ? noise_rows - 1 : row); // the host checked the range; never read outside
  const float *lg = logits + (size_t)i * V;
  const float *nz = noise + (size_t)row * V;
  float best = -__builtin_huge_valf();
  int bj = 0x7fffffff;
  for (int j = threadIdx.x; j < V; j += 256) {
    const float y = __fadd_rn(__fmul_rn(lg[j], inv_t), nz[j]);
    if (y > best || bj == 0x7fffffff) { // j grows, so on equal values the earlier index stays
      best = y;
      bj = j;
    }
  }
  sv[threadIdx.x] = best;
  si[threadIdx.x] = bj;
  __syncthreads();
  for (int h = 128; h >= 1; h >>= 1) {
    if (threadIdx.x < h) {
      const float ov = sv[threadIdx.x + h];
      const int oi = si[threadIdx.x + h];
      if (oi != 0x7fffffff && (si[threadIdx.x] == 0x7fffffff || ov > sv[threadIdx.x] ||
                               (ov == sv[threadIdx.x] && oi < si[threadIdx.x]))) {
        sv[threadIdx.x] = ov;
        si[threadIdx.x] = oi;
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) tokens[i] = si[0];
}

hipError_t launch_sample_tokens(const tr_ctx *c, const tr_kv *kv, const float *d_logits, const float *d_noise,
                                int32_t pos0, int32_t noise_rows, float inv_t, int32_t *d_tokens, hipStream_t st) {
  hipLaunchKernelGGL(k_sample_tokens, dim3(c->tree.n_nodes), dim3(256), 0, st, d_logits, d_noise, c->V, pos0, noise_rows,
                     inv_t, c->tree.depth, kv->d_len, d_tokens);
  return hipGetLastError();
}

hipError_t launch_accept_update(const tr_ctx *c, const tr_kv *kv, const int32_t *d_S, const int32_t *d_topk,
                                const int32_t *d_tokens, tr_step_out *d_out, hipStream_t st) {
  hipLaunchKernelGGL(k_accept_update, dim3(1), dim3(TR_MAX_NODES), 0, st, c->d_M, c->V, c->k, c->tree, d_S,
                     d_topk, d_tokens, kv->d_len, c->d_step_L, d_out, c->update_mode);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  const int blocks = kv->n_layers * kv->n_kv_heads;
  const size_t esz = dtype_size(kv->dtype);
  const size_t smem = 2 * (size_t)TR_MAX_LAYERS * kv->head_dim * esz;
  if (kv->dtype == TR_BF16)
    hipLaunchKernelGGL(k_compact_kv<bf16_t>, dim3(blocks), dim3(256), smem, st, (bf16_t *)kv->k, (bf16_t *)kv->v,
                       kv->capacity, kv->head_dim, kv->layout, c->d_step_L, d_out);
  else
    hipLaunchKernelGGL(k_compact_kv<float>, dim3(blocks), dim3(256), smem, st, (float *)kv->k, (float *)kv->v,
                       kv->capacity, kv->head_dim, kv->layout, c->d_step_L, d_out);
  return hipGetLastError();
}

// ---------------------------------------------------------------------------------------------
// Plain streaming kernels (measurement aids): a read-only pass and a copy over `slots` 16-byte slots,
// 256 workgroups of 512 threads, 4 independent nontemporal loads per thread in flight.
// ---------------------------------------------------------------------------------------------
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4s;
__global__ __launch_bounds__(512) void k_stream_read(const u32x4s *__restrict__ src, size_t slots, uint32_t *sink) {
  u32x4s acc = {0u, 0u, 0u, 0u};
  const size_t stride = (size_t)gridDim.x * 512;
  for (size_t i = (size_t)blockIdx.x * 512 + threadIdx.x; i < slots; i += 4 * stride) {
    u32x4s v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = i + u * stride < slots ? __builtin_nontemporal_load(src + i + u * stride) : u32x4s{0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < 4; ++u) acc ^= v[u];
  }
  if ((acc.x ^ acc.y ^ acc.z ^ acc.w) == 0x9E3779B9u && sink != nullptr) sink[0] = 1u; // keeps the loads alive
}
__global__ __launch_bounds__(512) void k_stream_copy(const u32x4s *__restrict__ src, u32x4s *__restrict__ dst, size_t slots) {
  const size_t stride = (size_t)gridDim.x * 512;
  for (size_t i = (size_t)blockIdx.x * 512 + threadIdx.x; i < slots; i += 4 * stride) {
    u32x4s v[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) v[u] = i + u * stride < slots ? __builtin_nontemporal_load(src + i + u * stride) : u32x4s{0u, 0u, 0u, 0u};
#pragma unroll
    for (int u = 0; u < 4; ++u)
      if (i + u * stride < slots) __builtin_nontemporal_store(v[u], dst + i + u * stride);
  }
}
hipError_t launch_stream(const void *src, void *dst, size_t bytes, hipStream_t st) {
  const size_t slots = bytes / 16;
  if (dst == nullptr)
    hipLaunchKernelGGL(k_stream_read, dim3(256), dim3(512), 0, st, (const u32x4s *)src, slots, (uint32_t *)nullptr);
  else
    hipLaunchKernelGGL(k_stream_copy, dim3(256), dim3(512), 0, st, (const u32x4s *)src, (u32x4s *)dst, slots);
  return hipGetLastError();
}

__global__ void k_advance_len(int32_t *d_len, int32_t by) { *d_len += by; }

hipError_t launch_advance_len(int32_t *d_len, int32_t by, hipStream_t st) {
  hipLaunchKernelGGL(k_advance_len, dim3(1), dim3(1), 0, st, d_len, by);
  return hipGetLastError();
}

} // namespace tr
