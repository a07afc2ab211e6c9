// Integer kernels of the Token Recycling step: draft-tree gather, per-row top-k, greedy accept,
// adjacency-matrix scatter and KV compaction.  All single-workgroup or tiny: the work is a few
// KB of dependent L2 accesses, so each kernel is shaped to be one launch with no host round trip.
#include <mutex>

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
    if (dep == d) { // a stored candidate outside [0, V) (a caller-made top-k buffer) is clamped like the root
      const int tk = M[(size_t)s[par] * k + rk];
      s[i] = tk < 0 ? 0 : (tk >= V ? V - 1 : tk);
    }
  }
  __syncthreads();
  if (live) S[i] = s[i];
}

hipError_t launch_build_tree(tr_ctx *c, const int32_t *d_root, int32_t *d_S, hipStream_t st) {
  return launch(k_build_tree, dim3(1), dim3(TR_MAX_NODES), 0, st, c->prof.next(PC_BUILD), c->d_M, c->V, c->k, c->tree,
                d_root, d_S);
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

// Two-stage variant for k <= 8, without workgroup barriers.  An element becomes one 64-bit key whose
// unsigned order is the total order of k_topk: the float mapped to an order-preserving unsigned (with
// -0 folded onto +0) in the high word, the complemented index in the low word; key 0 is "nothing".
// Stage 1: every wave owns TOPK_WAVE_ELEMS consecutive elements of a row, each lane holds 16 of them in
// registers together with their maximum, and k rounds of "wave-wide maximum, the owning lane drops it and
// recomputes its own" write the wave's k best keys.  Stage 2, one wave per row, merges the candidates of
// all waves of the row the same way (up to 16 per lane).
constexpr int TOPK_EPL = 16;                     // elements per lane
constexpr int TOPK_WAVE_ELEMS = 64 * TOPK_EPL;   // elements per stage-1 wave
constexpr int TOPK1_THREADS = 256;
constexpr int TOPK_MAX_WAVES_PER_ROW = 128;      // stage 2 holds 8 candidates per wave, 16 per lane

__device__ inline uint64_t topk_key(float v, int32_t idx) {
  uint32_t u = __float_as_uint(v + 0.0f); // -0 + 0 = +0
  u = (u & 0x80000000u) ? ~u : (u | 0x80000000u);
  return ((uint64_t)u << 32) | (uint32_t)~idx;
}
// Wave-wide maximum on the vector ALU alone: four data-parallel-primitive exchanges (lane ^ 1, lane ^ 2,
// mirror inside 8 lanes, mirror inside the row of 16) leave every lane with its row's maximum, and the
// four row maxima are read out as scalars.  All 64 lanes must be active.
template <int CTRL>
__device__ inline uint64_t dpp_u64(uint64_t x) {
  const uint32_t lo = (uint32_t)x, hi = (uint32_t)(x >> 32);
  const uint32_t l2 = (uint32_t)__builtin_amdgcn_update_dpp((int)lo, (int)lo, CTRL, 0xF, 0xF, false);
  const uint32_t h2 = (uint32_t)__builtin_amdgcn_update_dpp((int)hi, (int)hi, CTRL, 0xF, 0xF, false);
  return ((uint64_t)h2 << 32) | l2;
}
__device__ inline uint64_t readlane_u64(uint64_t x, int lane) {
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)x, lane);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readlane((int)(uint32_t)(x >> 32), lane);
  return ((uint64_t)hi << 32) | lo;
}
__device__ inline uint64_t max_u64(uint64_t a, uint64_t b) { return a > b ? a : b; }
__device__ inline uint64_t wave_max_u64(uint64_t x) {
  x = max_u64(x, dpp_u64<0xB1>(x));  // quad_perm [1,0,3,2]
  x = max_u64(x, dpp_u64<0x4E>(x));  // quad_perm [2,3,0,1]
  x = max_u64(x, dpp_u64<0x141>(x)); // row_half_mirror
  x = max_u64(x, dpp_u64<0x140>(x)); // row_mirror
  return max_u64(max_u64(readlane_u64(x, 0), readlane_u64(x, 16)), max_u64(readlane_u64(x, 32), readlane_u64(x, 48)));
}
// k rounds of maximum-with-replacement over the keys every lane holds; lane 0 writes the winners
__device__ inline void wave_select(uint64_t (&key)[TOPK_EPL], int32_t k, uint64_t *__restrict__ out) {
  uint64_t m = 0;
#pragma unroll
  for (int b = 0; b < TOPK_EPL; ++b) m = key[b] > m ? key[b] : m;
  for (int p = 0; p < k; ++p) {
    const uint64_t best = wave_max_u64(m);
    if ((threadIdx.x & 63) == 0) out[p] = best;
    if (m == best && best != 0) { // keys are unique (the index is part of them): one lane owns the winner
      m = 0;
#pragma unroll
      for (int b = 0; b < TOPK_EPL; ++b) {
        if (key[b] == best) key[b] = 0;
        m = key[b] > m ? key[b] : m;
      }
    }
  }
}

template <typename T>
__global__ __launch_bounds__(TOPK1_THREADS) void k_topk_stage1(const T *__restrict__ logits, int32_t V, int32_t k,
                                                                int32_t waves_per_row, uint64_t *__restrict__ cand) {
  const int rowi = blockIdx.y, lane = threadIdx.x & 63;
  const int w = blockIdx.x * (TOPK1_THREADS / 64) + (threadIdx.x >> 6); // wave index inside the row
  if (w >= waves_per_row) return;
  const T *row = logits + (size_t)rowi * V;
  const int lo = w * TOPK_WAVE_ELEMS;
  uint64_t key[TOPK_EPL];
#pragma unroll
  for (int b = 0; b < TOPK_EPL; ++b) {
    const int j = lo + b * 64 + lane;
    key[b] = j < V ? topk_key(to_f32<T>(row[j]), j) : 0;
  }
  wave_select(key, k, cand + ((size_t)rowi * waves_per_row + w) * 8);
}

__global__ __launch_bounds__(64) void k_topk_stage2(const uint64_t *__restrict__ cand, int32_t k, int32_t waves_per_row,
                                                    int32_t *__restrict__ out) {
  const int rowi = blockIdx.x, lane = threadIdx.x;
  const int n_cand = waves_per_row * 8; // slot c: wave c / 8, rank c % 8; ranks >= k were not written
  uint64_t key[TOPK_EPL];
#pragma unroll
  for (int b = 0; b < TOPK_EPL; ++b) {
    const int c = b * 64 + lane;
    key[b] = (c < n_cand && (c & 7) < k) ? cand[(size_t)rowi * n_cand + c] : 0;
  }
  __shared__ uint64_t win[8];
  wave_select(key, k, win);
  __syncthreads();
  if (lane < k) out[(size_t)rowi * k + lane] = (int32_t)~(uint32_t)win[lane];
}

hipError_t launch_topk(const void *logits, int32_t dtype, int32_t rows, int32_t V, int32_t k, int32_t *d_topk,
                       void *d_cand, Profiler *prof, hipStream_t st) {
  if (rows <= 0) return hipSuccess;
  const size_t esz = dtype_size(dtype);
  const int wpr = (V + TOPK_WAVE_ELEMS - 1) / TOPK_WAVE_ELEMS;
  if (k <= 8 && V >= 8 && wpr <= TOPK_MAX_WAVES_PER_ROW && d_cand != nullptr) {
    const int wg_per_row = (wpr + TOPK1_THREADS / 64 - 1) / (TOPK1_THREADS / 64);
    for (int r0 = 0; r0 < rows; r0 += TR_MAX_NODES) { // the candidate scratch holds TR_MAX_NODES rows
      const int nr = rows - r0 < TR_MAX_NODES ? rows - r0 : TR_MAX_NODES;
      const char *src = (const char *)logits + (size_t)r0 * V * esz;
      hipError_t e;
      if (dtype == TR_BF16)
        e = launch(k_topk_stage1<bf16_t>, dim3(wg_per_row, nr), dim3(TOPK1_THREADS), 0, st, prof_next(prof, PC_TOPK),
                   (const bf16_t *)src, V, k, wpr, (uint64_t *)d_cand);
      else
        e = launch(k_topk_stage1<float>, dim3(wg_per_row, nr), dim3(TOPK1_THREADS), 0, st, prof_next(prof, PC_TOPK),
                   (const float *)src, V, k, wpr, (uint64_t *)d_cand);
      if (e != hipSuccess) return e;
      e = launch(k_topk_stage2, dim3(nr), dim3(64), 0, st, prof_next(prof, PC_TOPK_MERGE), (const uint64_t *)d_cand, k,
                 wpr, d_topk + (size_t)r0 * k);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  }
  if (dtype == TR_BF16)
    return launch(k_topk<bf16_t>, dim3(rows), dim3(TOPK_THREADS), 0, st, prof_next(prof, PC_TOPK), (const bf16_t *)logits,
                  V, k, d_topk);
  return launch(k_topk<float>, dim3(rows), dim3(TOPK_THREADS), 0, st, prof_next(prof, PC_TOPK), (const float *)logits, V,
                k, d_topk);
}

size_t topk_scratch_bytes() { return (size_t)TR_MAX_NODES * TOPK_MAX_WAVES_PER_ROW * 8 * sizeof(uint64_t); }

// ---------------------------------------------------------------------------------------------
// argtopk without any allocation: the candidate scratch of the two-stage kernels is a file-scope device
// array (one copy per GPU, held until the process ends) instead of memory a context allocated.  In host
// code the array's name is only a stand-in: the address the kernels get comes from hipGetSymbolAddress,
// asked once per device with that device current.
// ---------------------------------------------------------------------------------------------
constexpr size_t TOPK_STATIC_BYTES = (size_t)TR_MAX_NODES * TOPK_MAX_WAVES_PER_ROW * 8 * sizeof(uint64_t); // 1 MiB
static __device__ __align__(256) unsigned char scratch[TOPK_STATIC_BYTES];

constexpr int MAX_DEVICES = 64;
static void *g_scratch_ptr[MAX_DEVICES];
static std::mutex g_scratch_mutex;

// Device address of this GPU's copy of `scratch`; nullptr (and *err set) if it cannot be had.
static void *static_scratch(hipError_t *err) {
  int dev = -1;
  *err = hipGetDevice(&dev);
  if (*err != hipSuccess) return nullptr;
  if (dev < 0 || dev >= MAX_DEVICES) {
    *err = hipErrorInvalidDevice;
    return nullptr;
  }
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (g_scratch_ptr[dev] == nullptr) {
    void *p = nullptr;
    *err = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (*err != hipSuccess || p == nullptr) {
      if (*err == hipSuccess) *err = hipErrorInvalidSymbol;
      return nullptr;
    }
    g_scratch_ptr[dev] = p;
  }
  return g_scratch_ptr[dev];
}

bool topk_static_fits(int32_t rows, int32_t V, int32_t k) {
  const int wpr = (V + TOPK_WAVE_ELEMS - 1) / TOPK_WAVE_ELEMS;
  return rows >= 0 && rows <= TR_MAX_NODES && V >= 8 && wpr <= TOPK_MAX_WAVES_PER_ROW && k >= 1 && k <= 8;
}

hipError_t launch_topk_static(const void *logits, int32_t dtype, int32_t rows, int32_t V, int32_t k, int32_t *d_topk,
                              hipStream_t st) {
  if (!topk_static_fits(rows, V, k)) return hipErrorInvalidValue;
  hipError_t e = hipSuccess;
  void *cand = static_scratch(&e);
  if (cand == nullptr) return e;
  // every candidate slot stage 2 reads is written by stage 1 of the same call, so nothing of the
  // previous call's contents needs clearing
  return launch_topk(logits, dtype, rows, V, k, d_topk, cand, nullptr, st);
}

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
  return launch(k_matrix_update, dim3(1), dim3(TR_MAX_NODES), 0, st, KernelTimer{}, c->d_M, c->V, c->k, c->tree.n_nodes,
                d_S, d_topk, c->update_mode);
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
  // everything that does not depend on the match is loaded up front, in one round trip
  const uint64_t anc0 = live ? t.anc[2 * i] : 0, anc1 = live ? t.anc[2 * i + 1] : 0;
  const int dep = live ? t.depth[i] : 0;
  const int par = live && i > 0 ? t.parent[i] : 0;
  const int L0 = i == 0 ? *d_len : 0;
  if (live) {
    int tk = S[i];
    sS[i] = tk < 0 ? 0 : (tk >= V ? V - 1 : tk);
    // the token the model emits at node i: its argmax, or the caller's draw under temperature sampling
    int ot = tokens != nullptr ? tokens[i] : topk[(size_t)i * k];
    sOut[i] = ot < 0 ? 0 : (ot >= V ? V - 1 : ot);
  }
  __syncthreads();
  const bool match = live && (i == 0 || sS[i] == sOut[par]);
  const uint64_t ballot = __ballot(match);
  if ((i & 63) == 0) mbits[i >> 6] = ballot;
  __syncthreads();
  if (live) {
    const bool ok = ((mbits[0] & anc0) == anc0) && ((mbits[1] & anc1) == anc1);
    if (ok) atomicMax(&best_key, dep * 256 + (255 - i));
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
    const int L = L0;
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

hipError_t launch_sample_tokens(tr_ctx *c, const tr_kv *kv, const float *d_logits, const float *d_noise,
                                int32_t pos0, int32_t noise_rows, float inv_t, int32_t *d_tokens, hipStream_t st) {
  return launch(k_sample_tokens, dim3(c->tree.n_nodes), dim3(256), 0, st, c->prof.next(PC_SAMPLE), d_logits, d_noise, c->V,
                pos0, noise_rows, inv_t, c->tree.depth, kv->d_len, d_tokens);
}

hipError_t launch_accept_update(tr_ctx *c, const tr_kv *kv, const int32_t *d_S, const int32_t *d_topk,
                                const int32_t *d_tokens, tr_step_out *d_out, hipStream_t st) {
  hipError_t e = launch(k_accept_update, dim3(1), dim3(TR_MAX_NODES), 0, st, c->prof.next(PC_ACCEPT), c->d_M, c->V, c->k,
                        c->tree, d_S, d_topk, d_tokens, kv->d_len, c->d_step_L, d_out, c->update_mode);
  if (e != hipSuccess) return e;
  const int blocks = kv->n_layers * kv->n_kv_heads;
  const size_t esz = dtype_size(kv->dtype);
  const size_t smem = 2 * (size_t)TR_MAX_LAYERS * kv->head_dim * esz;
  if (kv->dtype == TR_BF16)
    return launch(k_compact_kv<bf16_t>, dim3(blocks), dim3(256), smem, st, c->prof.next(PC_COMPACT), (bf16_t *)kv->k,
                  (bf16_t *)kv->v, kv->capacity, kv->head_dim, kv->layout, c->d_step_L, d_out);
  return launch(k_compact_kv<float>, dim3(blocks), dim3(256), smem, st, c->prof.next(PC_COMPACT), (float *)kv->k,
                (float *)kv->v, kv->capacity, kv->head_dim, kv->layout, c->d_step_L, d_out);
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
    return launch(k_stream_read, dim3(256), dim3(512), 0, st, KernelTimer{}, (const u32x4s *)src, slots, (uint32_t *)nullptr);
  return launch(k_stream_copy, dim3(256), dim3(512), 0, st, KernelTimer{}, (const u32x4s *)src, (u32x4s *)dst, slots);
}

__global__ void k_advance_len(int32_t *d_len, int32_t by) { *d_len += by; }

hipError_t launch_advance_len(int32_t *d_len, int32_t by, hipStream_t st) {
  return launch(k_advance_len, dim3(1), dim3(1), 0, st, KernelTimer{}, d_len, by);
}

} // namespace tr
