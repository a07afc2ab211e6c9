// Verification forward: one pass of a Llama-style decoder over the N tree nodes (Section 2.2).
// This file holds the orchestration and the shape-generic kernels (any head_dim, f32 or bf16
// storage, plain ALU arithmetic).  The bf16 hot shapes are routed to the MFMA kernels in
// tr_gemm_mfma.hip / tr_attn_mfma.hip.
//
// Arithmetic contract of the bf16 path (both generic and MFMA kernels): the residual stream, the
// softmax statistics, all accumulators and the logits are float32; operands of every contraction
// (normalised activations, rotated Q/K, V, attention output, SwiGLU output) are rounded to bf16.
#include "tr_internal.h"
#include "tr_kernels.h"

namespace tr {

static inline size_t align256(size_t x) { return (x + 255) & ~(size_t)255; }

Workspace plan_workspace(const tr_model &m) {
  Workspace w;
  const size_t esz = dtype_size(m.dtype);
  const size_t hq = (size_t)m.n_heads * m.head_dim, hk = (size_t)m.n_kv_heads * m.head_dim;
  size_t off = 0;
  auto take = [&](size_t bytes) { size_t o = off; off += align256(bytes); return o; };
  w.x = take((size_t)NP * m.d_model * 4);
  w.xn = take((size_t)NP * m.d_model * esz);
  w.qkv = take((size_t)NP * (hq + 2 * hk) * 4);
  w.q = take((size_t)NP * hq * esz);
  w.attn = take((size_t)NP * hq * esz);
  w.gu = take((size_t)NP * 2 * m.d_ffn * 4);
  w.h = take((size_t)NP * m.d_ffn * esz);
  w.rope = take((size_t)NP * m.head_dim * 4);
  w.logits = take((size_t)NP * m.vocab * 4);
  w.part_ml = take((size_t)ATTN_MAX_SPLITS * NP * m.n_heads * 2 * 4);
  w.part_acc = take((size_t)ATTN_MAX_SPLITS * NP * m.n_heads * m.head_dim * 4);
  w.total = off;
  return w;
}

// ---------------------------------------------------------------------------------------------
// Embedding gather + rotary table.  Row n: x[n,:] = E[tok[n],:]; cos/sin of (L + depth[n]) * f_i
// with f_i = theta^(-2i/hd), evaluated in double so that long positions keep float32 accuracy.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_embed_rope(const T *__restrict__ E, int32_t V, int32_t d,
                                                    const int32_t *__restrict__ tok, const int32_t *__restrict__ depth,
                                                    const int32_t *__restrict__ d_len, int32_t hd, float theta,
                                                    float *__restrict__ x, float *__restrict__ rope) {
  const int n = blockIdx.x;
  int t = tok[n];
  t = t < 0 ? 0 : (t >= V ? V - 1 : t);
  const T *src = E + (size_t)t * d;
  for (int j = threadIdx.x; j < d; j += blockDim.x) x[(size_t)n * d + j] = to_f32<T>(src[j]);
  const int half = hd / 2;
  const double pos = (double)(*d_len + depth[n]);
  for (int i = threadIdx.x; i < half; i += blockDim.x) {
    const double f = pow((double)theta, -2.0 * (double)i / (double)hd);
    double sn, cs;
    sincos(pos * f, &sn, &cs);
    rope[(size_t)n * hd + i] = (float)cs;
    rope[(size_t)n * hd + half + i] = (float)sn;
  }
}

// ---------------------------------------------------------------------------------------------
// RMSNorm: out[n,:] = T(x[n,:] * rsqrt(mean(x^2) + eps) * g)
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_rmsnorm(const float *__restrict__ x, const T *__restrict__ g, int32_t d,
                                                 float eps, T *__restrict__ out) {
  __shared__ float red[4];
  const int n = blockIdx.x;
  const float *row = x + (size_t)n * d;
  float ss = 0.f;
  for (int j = threadIdx.x; j < d; j += 256) {
    const float v = row[j];
    ss += v * v;
  }
  for (int off = 32; off > 0; off >>= 1) ss += __shfl_xor(ss, off);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = ss;
  __syncthreads();
  const float tot = (red[0] + red[1]) + (red[2] + red[3]);
  const float r = 1.0f / sqrtf(tot / (float)d + eps);
  for (int j = threadIdx.x; j < d; j += 256) out[(size_t)n * d + j] = from_f32<T>(row[j] * r * to_f32<T>(g[j]));
}

// ---------------------------------------------------------------------------------------------
// Generic linear: y[n,o] (+)= sum_k a[n,k] * w[o,k].  One wave per output feature and group of 16
// rows; lanes stride over k.  mode 0 = store, 1 = accumulate into y (residual add).
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_linear_generic(const T *__restrict__ a, const T *__restrict__ w, int32_t n,
                                                        int32_t K, int32_t O, float *__restrict__ y, int32_t ldy,
                                                        int32_t mode) {
  const int lane = threadIdx.x & 63;
  const int o = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int n0 = blockIdx.y * 16;
  if (o >= O) return;
  float acc[16];
#pragma unroll
  for (int j = 0; j < 16; ++j) acc[j] = 0.f;
  const T *wr = w + (size_t)o * K;
  for (int kk = lane; kk < K; kk += 64) {
    const float wv = to_f32<T>(wr[kk]);
#pragma unroll
    for (int j = 0; j < 16; ++j) {
      const int r = n0 + j;
      const float av = r < n ? to_f32<T>(a[(size_t)r * K + kk]) : 0.f;
      acc[j] += wv * av;
    }
  }
#pragma unroll
  for (int j = 0; j < 16; ++j) {
    float v = acc[j];
    for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off);
    acc[j] = v;
  }
  if (lane < 16 && n0 + lane < n) {
    float v = 0.f;
#pragma unroll
    for (int j = 0; j < 16; ++j)
      if (j == lane) v = acc[j];
    float *dst = y + (size_t)(n0 + lane) * ldy + o;
    *dst = mode ? (*dst + v) : v;
  }
}

template <typename T>
static hipError_t linear_generic(const void *a, const void *w, int32_t n, int32_t K, int32_t O, float *y, int32_t ldy,
                                 int32_t mode, hipStream_t st) {
  hipLaunchKernelGGL(k_linear_generic<T>, dim3((O + 3) / 4, (n + 15) / 16), dim3(256), 0, st, (const T *)a,
                     (const T *)w, n, K, O, y, ldy, mode);
  return hipGetLastError();
}

// h[n,f] = T(silu(g) * u) with gu = [gate | up], each F wide
template <typename T>
__global__ __launch_bounds__(256) void k_swiglu(const float *__restrict__ gu, int32_t F, T *__restrict__ h) {
  const int n = blockIdx.y;
  const int f = blockIdx.x * 256 + threadIdx.x;
  if (f >= F) return;
  const float g = gu[(size_t)n * 2 * F + f], u = gu[(size_t)n * 2 * F + F + f];
  h[(size_t)n * F + f] = from_f32<T>(g / (1.0f + expf(-g)) * u);
}

// ---------------------------------------------------------------------------------------------
// Rotary embedding + KV write.  Block (n, head) over the concatenated [q heads | k heads | v heads].
// Rotated q -> q[n, h, :]; rotated k -> K[layer][h][L+n][:]; v -> V[layer][h][:][L+n].
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(128) void k_rope_kv(const float *__restrict__ qkv, const float *__restrict__ rope,
                                                 int32_t H, int32_t Hkv, int32_t hd, int32_t cap,
                                                 const int32_t *__restrict__ d_len, T *__restrict__ q,
                                                 T *__restrict__ Kl, T *__restrict__ Vl) {
  const int n = blockIdx.x, hh = blockIdx.y;
  const int half = hd / 2;
  const int width = (H + 2 * Hkv) * hd;
  const float *src = qkv + (size_t)n * width + (size_t)hh * hd;
  const int pos = *d_len + n;
  if (hh < H + Hkv) {
    for (int i = threadIdx.x; i < half; i += blockDim.x) {
      const float c = rope[(size_t)n * hd + i], s = rope[(size_t)n * hd + half + i];
      const float a = src[i], b = src[i + half];
      const T ra = from_f32<T>(a * c - b * s), rb = from_f32<T>(b * c + a * s);
      if (hh < H) {
        T *dst = q + ((size_t)n * H + hh) * hd;
        dst[i] = ra;
        dst[i + half] = rb;
      } else {
        T *dst = Kl + ((size_t)(hh - H) * cap + pos) * hd;
        dst[i] = ra;
        dst[i + half] = rb;
      }
    }
  } else {
    T *dst = Vl + (size_t)(hh - H - Hkv) * hd * cap + pos;
    for (int i = threadIdx.x; i < hd; i += blockDim.x) dst[(size_t)i * cap] = from_f32<T>(src[i]);
  }
}

// ---------------------------------------------------------------------------------------------
// Generic tree attention (Section 2.2 "Tree Attention"): block (node n, head h).  Keys are the
// committed positions 0..L-1 and the tree nodes j whose bit is set in anc[n] (cache position L+j);
// everything else is skipped exactly.  Online softmax over chunks of 256 keys.
// ---------------------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_attn_generic(const T *__restrict__ q, const T *__restrict__ Kl,
                                                      const T *__restrict__ Vl, int32_t H, int32_t Hkv, int32_t hd,
                                                      int32_t cap, int32_t n_nodes, const uint64_t *__restrict__ anc,
                                                      const int32_t *__restrict__ d_len, T *__restrict__ out) {
  __shared__ float sq[256];
  __shared__ float sp[256];
  __shared__ float red[4];
  const int n = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
  const int hk = h / (H / Hkv);
  const int L = *d_len;
  const uint64_t a0 = anc[2 * n], a1 = anc[2 * n + 1];
  const T *Kh = Kl + (size_t)hk * cap * hd;
  const T *Vh = Vl + (size_t)hk * hd * cap;
  if (tid < hd) sq[tid] = to_f32<T>(q[((size_t)n * H + h) * hd + tid]);
  __syncthreads();
  const float scale = 1.0f / sqrtf((float)hd);
  float m = -1e30f, l = 0.f, acc = 0.f; // acc: output element tid (< hd)
  const int total = L + n_nodes;
  for (int base = 0; base < total; base += 256) {
    const int j = base + tid;
    bool vis = j < L;
    if (!vis && j < total) {
      const int t = j - L;
      vis = t < 64 ? ((a0 >> t) & 1) : ((a1 >> (t - 64)) & 1);
    }
    float s = -1e30f;
    if (vis) {
      const T *kr = Kh + (size_t)j * hd;
      float dot = 0.f;
      for (int e = 0; e < hd; ++e) dot += sq[e] * to_f32<T>(kr[e]);
      s = dot * scale;
    }
    float cm = s;
    for (int off = 32; off > 0; off >>= 1) cm = fmaxf(cm, __shfl_xor(cm, off));
    if ((tid & 63) == 0) red[tid >> 6] = cm;
    __syncthreads();
    cm = fmaxf(fmaxf(red[0], red[1]), fmaxf(red[2], red[3]));
    const float m_new = fmaxf(m, cm);
    const float p = vis ? expf(s - m_new) : 0.f;
    sp[tid] = p;
    float ps = p;
    for (int off = 32; off > 0; off >>= 1) ps += __shfl_xor(ps, off);
    __syncthreads(); // red (max) consumed by everyone, sp complete
    if ((tid & 63) == 0) red[tid >> 6] = ps;
    __syncthreads();
    const float corr = expf(m - m_new);
    l = l * corr + ((red[0] + red[1]) + (red[2] + red[3]));
    m = m_new;
    if (tid < hd) {
      acc *= corr;
      const T *vr = Vh + (size_t)tid * cap + base;
      const int cnt = total - base < 256 ? total - base : 256;
      for (int e = 0; e < cnt; ++e) {
        const float pe = sp[e];
        if (pe != 0.f) acc += pe * to_f32<T>(vr[e]);
      }
    }
    __syncthreads();
  }
  if (tid < hd) out[((size_t)n * H + h) * hd + tid] = from_f32<T>(acc / l);
}

// ---------------------------------------------------------------------------------------------
// orchestration
// ---------------------------------------------------------------------------------------------
#define TR_TRY(expr)                   \
  do {                                 \
    hipError_t e__ = (expr);           \
    if (e__ != hipSuccess) return e__; \
  } while (0)

template <typename T>
static hipError_t attention_dispatch(const tr_kv &kv, int32_t layer, int32_t H, const TreeDev &tree, int32_t n,
                                     const T *q, T *out, const Workspace *w, unsigned char *ws, hipStream_t st) {
  const size_t lsz = (size_t)kv.n_kv_heads * kv.capacity * kv.head_dim;
  const T *Kl = (const T *)kv.k + (size_t)layer * lsz;
  const T *Vl = (const T *)kv.v + (size_t)layer * lsz;
  if (sizeof(T) == 2 && attn_mfma_supported(kv.head_dim, n) && w != nullptr) {
    return launch_attn_mfma((const bf16_t *)q, (const bf16_t *)Kl, (const bf16_t *)Vl, H, kv.n_kv_heads, kv.capacity,
                            n, tree.anc, kv.d_len, kv.len_bound + n, (float *)(ws + w->part_ml),
                            (float *)(ws + w->part_acc), (bf16_t *)out, st);
  }
  hipLaunchKernelGGL(k_attn_generic<T>, dim3(n, H), dim3(256), 0, st, q, Kl, Vl, H, kv.n_kv_heads, kv.head_dim,
                     kv.capacity, n, tree.anc, kv.d_len, out);
  return hipGetLastError();
}

template <typename T>
static hipError_t linear_dispatch(const T *a, const T *w, int32_t n, int32_t K, int32_t O, float *y, int32_t ldy,
                                  int32_t mode, hipStream_t st) {
  if (sizeof(T) == 2 && gemm_mfma_supported(n, K, O))
    return launch_gemm_mfma((const bf16_t *)a, (const bf16_t *)w, nullptr, n, K, O, y, ldy,
                            mode ? GEMM_ADD : GEMM_STORE, nullptr, st);
  return linear_generic<T>(a, w, n, K, O, y, ldy, mode, st);
}

template <typename T>
static hipError_t forward_t(const tr_model &m, const tr_kv &kv, const TreeDev &tree, int32_t n, const int32_t *tok,
                            float *logits_out, unsigned char *ws, hipStream_t st) {
  const Workspace w = plan_workspace(m);
  const int d = m.d_model, H = m.n_heads, Hkv = m.n_kv_heads, hd = m.head_dim, F = m.d_ffn;
  const int hq = H * hd, hk = Hkv * hd, wq = hq + 2 * hk;
  float *x = (float *)(ws + w.x);
  T *xn = (T *)(ws + w.xn);
  float *qkv = (float *)(ws + w.qkv);
  T *q = (T *)(ws + w.q);
  T *attn = (T *)(ws + w.attn);
  float *gu = (float *)(ws + w.gu);
  T *hbuf = (T *)(ws + w.h);
  float *rope = (float *)(ws + w.rope);
  const size_t lsz = (size_t)Hkv * kv.capacity * hd;

  hipLaunchKernelGGL(k_embed_rope<T>, dim3(n), dim3(256), 0, st, (const T *)m.embed, m.vocab, d, tok, tree.depth,
                     kv.d_len, hd, m.rope_theta, x, rope);
  TR_TRY(hipGetLastError());
  for (int l = 0; l < m.n_layers; ++l) {
    const tr_layer &lw = m.layers[l];
    hipLaunchKernelGGL(k_rmsnorm<T>, dim3(n), dim3(256), 0, st, x, (const T *)lw.attn_norm, d, m.rms_eps, xn);
    TR_TRY(hipGetLastError());
    TR_TRY(linear_dispatch<T>(xn, (const T *)lw.wq, n, d, hq, qkv, wq, 0, st));
    TR_TRY(linear_dispatch<T>(xn, (const T *)lw.wk, n, d, hk, qkv + hq, wq, 0, st));
    TR_TRY(linear_dispatch<T>(xn, (const T *)lw.wv, n, d, hk, qkv + hq + hk, wq, 0, st));
    hipLaunchKernelGGL(k_rope_kv<T>, dim3(n, H + 2 * Hkv), dim3(128), 0, st, qkv, rope, H, Hkv, hd, kv.capacity,
                       kv.d_len, q, (T *)kv.k + (size_t)l * lsz, (T *)kv.v + (size_t)l * lsz);
    TR_TRY(hipGetLastError());
    TR_TRY(attention_dispatch<T>(kv, l, H, tree, n, q, attn, &w, ws, st));
    TR_TRY(linear_dispatch<T>(attn, (const T *)lw.wo, n, hq, d, x, d, 1, st));
    hipLaunchKernelGGL(k_rmsnorm<T>, dim3(n), dim3(256), 0, st, x, (const T *)lw.ffn_norm, d, m.rms_eps, xn);
    TR_TRY(hipGetLastError());
    if (sizeof(T) == 2 && gemm_mfma_supported(n, d, F)) {
      TR_TRY(launch_gemm_mfma((const bf16_t *)xn, (const bf16_t *)lw.w_gate, (const bf16_t *)lw.w_up, n, d, F, nullptr,
                              F, GEMM_SWIGLU, (bf16_t *)hbuf, st));
    } else {
      TR_TRY(linear_generic<T>(xn, lw.w_gate, n, d, F, gu, 2 * F, 0, st));
      TR_TRY(linear_generic<T>(xn, lw.w_up, n, d, F, gu + F, 2 * F, 0, st));
      hipLaunchKernelGGL(k_swiglu<T>, dim3((F + 255) / 256, n), dim3(256), 0, st, gu, F, hbuf);
      TR_TRY(hipGetLastError());
    }
    TR_TRY(linear_dispatch<T>(hbuf, (const T *)lw.w_down, n, F, d, x, d, 1, st));
  }
  if (logits_out != nullptr) {
    hipLaunchKernelGGL(k_rmsnorm<T>, dim3(n), dim3(256), 0, st, x, (const T *)m.final_norm, d, m.rms_eps, xn);
    TR_TRY(hipGetLastError());
    TR_TRY(linear_dispatch<T>(xn, (const T *)m.lm_head, n, d, m.vocab, logits_out, m.vocab, 0, st));
  }
  return hipSuccess;
}

hipError_t run_forward(const tr_model &m, const tr_kv &kv, const TreeDev &tree, int32_t n, const int32_t *d_tokens,
                       float *write_logits, void *ws, hipStream_t st) {
  if (m.dtype == TR_BF16) return forward_t<bf16_t>(m, kv, tree, n, d_tokens, write_logits, (unsigned char *)ws, st);
  return forward_t<float>(m, kv, tree, n, d_tokens, write_logits, (unsigned char *)ws, st);
}

hipError_t run_tree_attention(const tr_kv &kv, int32_t layer, int32_t H, const TreeDev &tree, const void *d_q,
                              void *d_out, void *ws, hipStream_t st) {
  // standalone op: the split partials sit at the start of the caller's workspace
  Workspace w;
  w.part_ml = 0;
  w.part_acc = align256((size_t)ATTN_MAX_SPLITS * NP * H * 2 * 4);
  if (kv.dtype == TR_BF16)
    return attention_dispatch<bf16_t>(kv, layer, H, tree, tree.n_nodes, (const bf16_t *)d_q, (bf16_t *)d_out, &w,
                                      (unsigned char *)ws, st);
  return attention_dispatch<float>(kv, layer, H, tree, tree.n_nodes, (const float *)d_q, (float *)d_out, nullptr,
                                   (unsigned char *)ws, st);
}

hipError_t run_linear(const void *x, const void *w, int32_t dtype, int32_t n, int32_t in_f, int32_t out_f, float *y,
                      hipStream_t st) {
  if (dtype == TR_BF16) return linear_dispatch<bf16_t>((const bf16_t *)x, (const bf16_t *)w, n, in_f, out_f, y, out_f, 0, st);
  return linear_dispatch<float>((const float *)x, (const float *)w, n, in_f, out_f, y, out_f, 0, st);
}

} // namespace tr
